"""MI355X-native OIM + SPU token compression (hand-written HIP behind a C ABI).

``workloads`` holds the seeded input generators; ``binding`` the ctypes layer over ``libluvc.so``.
"""
