"""MI355X-native layout-elided transformer chains (SmartMem, arxiv 2404.13528).

Importing this package loads nothing; `paper_2404_13528_amd.binding` loads the
HIP library on first use and raises if it is missing.
"""
