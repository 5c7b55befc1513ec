"""MI355X-native staged multi-tenant CNN inference (arXiv 2111.14255): Python side of libmtsched.so."""
import os as _os


def _runtime_environment():
    """Settings the HIP runtime reads when it initialises (the first HIP call of the process), so they are made on
    import of the package, before anything touches the GPU.

    GPU_MAX_HW_QUEUES: hardware queues the runtime shares among the plain streams of the process.  With the HIP
    default of 4 the streams of three tenants and the main stream share queues with each other and with the
    framework's own streams, and concurrent tenants then serialise (measured on MI355X, ResNet-18 + VGG-16 +
    MobileNetV2 all concurrent on plain streams: 0.54 ms with 4 queues, 0.42 ms with 8 or 16; with one issuing thread
    per stream 0.56 against 0.36 ms).  Raised to 8 if lower; a larger value already set is kept; MTSCHED_HW_QUEUES=<n>
    (1..32) forces a value, for measurements.  The price: with more than 4 queues the replay of some captured
    multi-stage schedules is slow in one of the two capture orders (1 to 2.7 ms instead of 0.4 to 0.6 ms), which is
    why the library captures a schedule in both orders and keeps the faster graph.
    HIP_FORCE_DEV_KERNARG: kernel arguments in device memory; in host memory every launch starts with a read over
    the host link (848 against 578 us for the 98 launches of that pass).  The runtime of this image already defaults
    to it; set here so that another default does not change the numbers.
    HSA_ENABLE_INTERRUPT=0: host waits for device signals (hipEventSynchronize at the end of a run and in host-side
    stage barriers) poll the signal instead of sleeping until the driver's interrupt wakes the thread.  Measured on
    MI355X: the same three-tenant pass 0.294 -> 0.286 ms per step on the host's clock (makespan 0.279 -> 0.272 ms),
    even two- to seven-stage schedules 4 to 8 % shorter.  The price is a busy host thread per waiting call; a value
    already set in the environment is kept.

    MTSCHED_KEEP_ENV=1 switches all of this off: the process environment is left as it is (for hosts that set these
    variables themselves, or that must not have a polling thread).  None of the settings has any effect when the HIP
    runtime was initialised before this package is imported."""
    if _os.environ.get("MTSCHED_KEEP_ENV", "") not in ("", "0"):
        return
    want = _os.environ.get("MTSCHED_HW_QUEUES")
    try:
        have = int(_os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0)
    except ValueError:
        have = 0
    if want:
        _os.environ["GPU_MAX_HW_QUEUES"] = str(max(1, min(32, int(want))))
    elif have < 8:
        _os.environ["GPU_MAX_HW_QUEUES"] = "8"
    _os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")
    _os.environ.setdefault("HSA_ENABLE_INTERRUPT", "0")


_runtime_environment()

from . import binding  # noqa: E402,F401
