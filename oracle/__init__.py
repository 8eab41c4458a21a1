"""CPU oracle of Dual-scope attention: TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this
package; it shares no code with paper_2406_16260_amd and never imports it.
"""
