"""What the measurements ran on: ROCm/HIP version, device, partition modes, memory clock.

Partition modes and clocks come from `rocm-smi --json`, run as a child process; call `environment()`
before the process touches the GPU.  Under a profiler (which preloads its own library into every
child) the tool is not run and those fields are None.
"""
import json
import os
import subprocess
from typing import Dict, Optional


def _smi() -> Optional[Dict[str, str]]:
    if any("rocprof" in v.lower() for v in (os.environ.get("LD_PRELOAD", ""), os.environ.get("ROCP_TOOL_LIBRARIES", ""))):
        return None
    try:
        out = subprocess.run(["rocm-smi", "--showcomputepartition", "--showmemorypartition", "--showclocks", "--json"],
                             capture_output=True, text=True, timeout=30)
        cards = json.loads(out.stdout)
        return next(iter(cards.values())) if cards else None
    except (OSError, ValueError, subprocess.SubprocessError):
        return None


def environment() -> Dict[str, Optional[str]]:
    """Static facts only (no GPU call is made here apart from what `rocm-smi` does in its own process)."""
    card = _smi() or {}
    import torch
    try:
        with open("/opt/rocm/.info/version") as f:
            rocm = f.read().strip()
    except OSError:
        rocm = None
    return {"rocm": rocm, "torch_hip": getattr(torch.version, "hip", None), "torch": torch.__version__,
            "compute_partition": card.get("Compute Partition"), "memory_partition": card.get("Memory Partition"),
            "mclk": (card.get("mclk clock speed:") or "").strip("()") or None}


def device_facts() -> Dict[str, object]:
    """Name, architecture, CU count and memory of device 0 (initialises the GPU)."""
    import torch
    p = torch.cuda.get_device_properties(0)
    return {"device": p.name, "arch": getattr(p, "gcnArchName", None), "compute_units": p.multi_processor_count,
            "memory_gib": round(p.total_memory / (1 << 30), 2)}
