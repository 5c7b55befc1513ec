"""placeholder; replaced below"""
def speedup(sequential_ms, ours_ms):
    return sequential_ms / ours_ms
