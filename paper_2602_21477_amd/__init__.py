"""MI355X-native IVF search / insert hot path behind a C-ABI library (libpancake).

``workload`` generates the seeded synthetic inputs; ``binding`` wraps the C-ABI
entry points (``pk_index_build``, ``pk_insert``, ``pk_search`` ...) one to one.
"""
