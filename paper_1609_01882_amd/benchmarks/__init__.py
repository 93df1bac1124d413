"""Timing scripts for the workloads other than the headline one (which bench.py at the repository
root measures): the 128-bit flat scan, the inverted-file batch search and the k-NN-graph mode.
Each builds its index with the library, runs the search on cuda:0 and prints one JSON line.

    python -m paper_1609_01882_amd.benchmarks.flat128
    python -m paper_1609_01882_amd.benchmarks.ivf
    python -m paper_1609_01882_amd.benchmarks.graph
"""
