"""Block programs, substitution rules and the fusion algorithm of "Blockbuster,
Part 1" as a host-side tool: derives the fused loop nests the HIP kernels of
this package implement (Examples 1-3) from the array programs."""
from .algorithm import PRIORITY, extend_once, fuse, fuse_in_place, saturate, saturate_all  # noqa: F401
from .emit import intermediate_buffers, listing, nest, skeleton  # noqa: F401
from .lower import EXAMPLES, Program, example1, example2, example3  # noqa: F401
