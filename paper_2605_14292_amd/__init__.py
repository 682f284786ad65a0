"""MI355X-native retention step of the alpha selector (score -> greedy
V-diversity selection -> K/V compaction) behind a C-ABI HIP library."""
