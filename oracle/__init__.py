"""fp64 CPU oracle of the PreFT adapter-apply path -- test infrastructure, never product code."""
