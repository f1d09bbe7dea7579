"""Random cache-line read benchmark for MI355X (gfx950): HIP library + thin binding.

Implements the benchmark, window placement and pair probe of "Enabling full-speed
random access to the entire memory on the A100 GPU" (Sec. 2.1-2.4) for CDNA4.
"""
from .binding import (BCAST_DEFAULT, BCAST_DPP, BCAST_LDS, BCAST_READLANE, MODE_AUTO, MODE_FLAT,
                      MODE_TICKET, MODE_STREAM, SPLIT_DEFAULT, SPLIT_ON, SPLIT_OFF, NT_DEFAULT, NT_OFF, NT_ON, RR_CU_EXCLUDED, RR_EHIP, RR_EINVAL, RR_EPLACE, RR_OK, RandlineError,
                      ReadResult, WindowMap, enumerate_cus, fill, groups_from_heatmap, lib, library_path,
                      probe_cus, probe_pair, rand_read, rand_read_noalloc, rand_read_batch, ReadBatch, rand_update, OP_ADD, OP_WRITE, seq_read, copy, chase, shutdown,
                      Region, region_create, region_granularity, zones_from_pair_rates, detect_zones, ZONE_NO_WARMUP, last_kernel, describe_read)

__all__ = ["BCAST_DEFAULT", "BCAST_DPP", "BCAST_LDS", "BCAST_READLANE", "MODE_AUTO", "MODE_FLAT",
           "MODE_TICKET", "MODE_STREAM", "SPLIT_DEFAULT", "SPLIT_ON", "SPLIT_OFF", "NT_DEFAULT", "NT_OFF", "NT_ON", "RR_CU_EXCLUDED", "RR_EHIP", "RR_EINVAL", "RR_EPLACE", "RR_OK", "RandlineError",
           "ReadResult", "WindowMap", "enumerate_cus", "fill", "groups_from_heatmap", "lib",
           "library_path", "probe_cus", "probe_pair", "rand_read", "rand_read_noalloc", "rand_read_batch", "ReadBatch", "seq_read", "copy", "chase", "rand_update", "OP_ADD", "OP_WRITE", "shutdown",
           "Region", "region_create", "region_granularity", "zones_from_pair_rates", "detect_zones", "ZONE_NO_WARMUP", "last_kernel", "describe_read"]
