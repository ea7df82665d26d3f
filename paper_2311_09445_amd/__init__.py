"""MI355X-native prioritized replay buffer (K-ary sum tree) behind a C-ABI.

``workloads`` (seeded synthetic inputs) is importable without the HIP library;
the binding in ``per`` loads ``libper_hip.so`` on first use and fails loudly if
it has not been built.
"""
