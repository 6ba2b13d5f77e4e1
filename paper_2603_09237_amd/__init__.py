"""MI355X-native hot path of MORLAX (preference-conditioned rollout-and-update step).

Sub-modules: `configs` (workload shapes), `inputs` (seeded synthetic tensors),
`binding` (ctypes view of the C-ABI library built from `csrc/`).  Importing the
package loads nothing native; `binding.load()` does and fails loudly if the
library has not been built.
"""
