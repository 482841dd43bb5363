"""MI355X-native shard path of the column-partitioned word2vec parameter server (arXiv 1606.08495).

``paper_1606_08495_amd.w2v`` is the thin binding over the C-ABI library (libw2v_shard.so, built
from csrc/ for gfx950); ``paper_1606_08495_amd.workloads`` makes seeded synthetic inputs.
Importing the package loads nothing; the library is opened on first use and a missing library is
an error, never a fallback.
"""
