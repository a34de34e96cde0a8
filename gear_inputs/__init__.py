"""Seeded synthetic inputs for the Gear Training sparse-part step.

This package only *draws inputs* (workload shapes, page-view batches, id
distributions).  It holds none of the method's arithmetic and imports neither
the CPU oracle nor the HIP library, so both can be fed from it.
"""
from .configs import GearWorkload, WORKLOADS, get_workload  # noqa: F401
from .pageviews import PageViewBatch, PageViewSource, ZipfIds  # noqa: F401
