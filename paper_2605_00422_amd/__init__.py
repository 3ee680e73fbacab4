"""MI355X-native W1A6 quantized linear forward of BWLA (arxiv 2605.00422).

`paper_2605_00422_amd.binding` is the ctypes binding over the C-ABI library in `csrc/`;
`paper_2605_00422_amd.inputs` draws the seeded synthetic layers.  Nothing is loaded at
package import time.
"""
