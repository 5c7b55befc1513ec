"""MI355X-native staged multi-tenant CNN inference (arXiv 2111.14255): Python side of libmtsched.so."""
import os as _os


def _runtime_environment():
    """Settings the HIP runtime reads when it initialises (the first HIP call of the process), so they are made on
    import of the package, before anything touches the GPU.

    HIP_FORCE_DEV_KERNARG: kernel arguments in device memory; in host memory every launch starts with a read over
    the host link (measured on MI355X: 848 against 578 us for the 98 launches of the ResNet-18 + VGG-16 +
    MobileNetV2 pass).  The runtime of this image already defaults to it; set here so that another default does not
    change the numbers.
    GPU_MAX_HW_QUEUES is left as the environment has it (the HIP default is 4): every tenant stream is created with a
    CU mask and therefore owns a hardware queue whatever that number is.  MTSCHED_HW_QUEUES=<n> (1..32) sets it, for
    measurements only: with more than 4 queues the replay of some captured multi-stage schedules took 1 to 2.7 ms
    instead of 0.4 to 0.6 ms."""
    want = _os.environ.get("MTSCHED_HW_QUEUES")
    if want:
        _os.environ["GPU_MAX_HW_QUEUES"] = str(max(1, min(32, int(want))))
    _os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")


_runtime_environment()

from . import binding  # noqa: E402,F401
