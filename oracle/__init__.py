"""CPU oracle for the SVG-EAR attention hot path -- test infrastructure only.

Importable from tests/, the smoke check and the benchmark's cpu_baseline leg; the product
package never imports it.
"""
from . import svgear_oracle  # noqa: F401
